"""MI355X-native paged sparse attention (forward + backward) for OOMB-style
chunk-recurrent long-context training.  See `api` for the Python binding of the
C-ABI library and `workloads` for the seeded synthetic inputs."""
