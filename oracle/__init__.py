"""CPU oracle of the TT-EmbeddingBag path: test infrastructure, not product code."""
