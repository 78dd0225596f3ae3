"""HashEvict's pre-attention KV-cache eviction path for AMD MI355X (gfx950).

``binding``  ctypes binding of the C-ABI HIP library (``include/lshe.h``)
``state``    device buffers of a fixed-budget cache (allocation + calls into ``binding``)
``synth``    seeded synthetic workloads (no method arithmetic)
``build``    compiles ``csrc/`` into ``liblshe.so`` with hipcc

Importing the package does not load the library; the first call into ``binding`` does,
and raises if it has not been built.
"""
