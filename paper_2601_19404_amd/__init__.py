"""MI355X-native suffix-rollout hot path of RPO (arXiv 2601.19404): a HIP library
behind a C ABI (include/rpo.h) plus this thin ctypes binding."""
