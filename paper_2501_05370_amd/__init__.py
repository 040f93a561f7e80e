"""MI355X-native speculative sampling for diffusion chains: HIP library + thin ctypes binding.

``binding`` forwards to the C entry points of ``include/sd.h`` / ``include/sdden.h``;
``sampler`` holds the host-side window loop; ``build`` compiles the library in-tree.
Nothing here computes on the CPU: without the built library the binding raises.
"""
