"""MI355X implementation of AMPNet's asynchronous model-parallel training
hot path (arXiv 1705.09786): a persistent HIP kernel behind a C boundary
(include/amp.h), with a thin ctypes binding in `binding`."""
