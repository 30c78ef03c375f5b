"""MI355X-native executor for SCCL-style collective schedules (one GPU, P virtual ranks).

Submodules
  sccl           ctypes binding of the C-ABI library (csrc/, include/sccl.h)
  schedule_file  reader for the text schedule files under schedules/
  inputs         seeded synthetic rank buffers (no method arithmetic)
"""
