"""TEST INFRASTRUCTURE ONLY: slow, plain CPU definitions used to check the GPU library.

Nothing in the product package imports this; only tests, the smoke check and the
benchmark's cpu_baseline leg do.  It shares no code with the HIP path.

  direct     conv2d by its definition (C, int32 accumulation)        -- pinned
  layouts    pack / weight-pack / im2col index maps, GEMM unit (numpy) -- pinned
  selection  candidate-selection overheads O_MAC, O_Data (Sec. 4.4)   -- pinned
"""
