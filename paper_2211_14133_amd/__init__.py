"""MI355X-native K-FAC work items (curvature, inversion, precondition) behind a C ABI."""
