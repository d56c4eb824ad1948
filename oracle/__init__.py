"""CPU oracle for the PEQA quantized linear layer -- test infrastructure only."""
