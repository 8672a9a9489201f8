"""CPU oracle of the FFT-sparsifying gradient codec: test infrastructure only."""
