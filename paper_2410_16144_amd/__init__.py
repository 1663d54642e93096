"""MI355X (gfx950) BitLinear library for the ternary kernels of arXiv 2410.16144.

  binding  -- ctypes mirror of include/bitlinear.h (raw pointers in, status checked)
  ops      -- torch-tensor conveniences over the binding (allocation + current stream only)
  synth    -- seeded synthetic inputs and the paper's model shapes
  build    -- compiles csrc/*.hip into libbitlinear.so with hipcc

All arithmetic runs in the HIP kernels under csrc/.  Nothing here falls back to the CPU.
"""
