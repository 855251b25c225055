"""MI355X-native hot path of Dynamic Expert Sharing: one MoE layer over a
parallel-decoding block.  The compute lives in the C-ABI library built from
`csrc/` (see `include/des.h`); `binding` marshals arguments to it and
`workloads` draws the seeded synthetic inputs.  Nothing is imported eagerly so
that `workloads` can be used without the compiled library."""
__all__ = ["binding", "workloads"]
