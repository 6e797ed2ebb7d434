"""CPU oracle (test infrastructure only).  See decoder_layer.py for the contract."""
