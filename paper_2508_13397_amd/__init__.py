"""MI355X-native emulated lane-aware all-reduce (segmented k-way reduce schedules on one GPU)."""
