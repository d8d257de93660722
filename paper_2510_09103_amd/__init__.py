"""AdaPM optimizer step for AMD MI355X: C-ABI HIP library + thin ctypes binding."""
