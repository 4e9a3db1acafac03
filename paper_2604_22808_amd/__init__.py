"""freqattn: FreqFormer's frequency-domain heterogeneous attention for one MI355X (HIP library + ctypes binding)."""
