"""MI355X-native waveform -> spectrogram transforms (STFT, Mel, CQT) behind a C ABI.

``signals`` (input generators) can be imported on its own; the GPU binding is
loaded lazily by ``paper_1912_12055_amd.binding``.
"""
