"""CPU oracle for the KNN-SSD decode path: test infrastructure, never imported by the product."""
